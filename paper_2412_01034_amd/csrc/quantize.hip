// Round-to-nearest quantisers and (un)packers (Sec. 2.1 RTN; Sec. 5.1 4-bit formats).
//
// These are one-off, HBM-bound elementwise/reduction kernels; what matters is
// that the codes are bit-identical to the definition: fp32 arithmetic with
// correctly rounded division (compile with -fhip-fp32-correctly-rounded-divide-sqrt,
// no fast-math) and rint = ties-to-even.
#include "qail_internal.h"

namespace qail {

namespace {

constexpr int kQuantBlock = 256;

// Smallest fp16 >= v, for finite 0 <= v <= 65504, as a bit pattern.
__device__ __forceinline__ uint16_t f32_to_f16_bits_up(float v) {
    _Float16 h = (_Float16)v;  // nearest even
    uint16_t b = __builtin_bit_cast(uint16_t, h);
    if ((float)h < v) b += 1;  // positive fp16 patterns are ordered like integers
    return b;
}

__device__ __forceinline__ void load8(const float* p, float (&v)[8]) {
    const float4 a = *reinterpret_cast<const float4*>(p);
    const float4 b = *reinterpret_cast<const float4*>(p + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
    v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}

// One block per row.  A team of LPG lanes (power of two) owns one group at a
// time; lane t of the team covers 8-element words t, t+LPG, ... of the group.
template <int LPG>
__global__ __launch_bounds__(kQuantBlock) void quantize_asym_kernel(
    const float* __restrict__ w, uint32_t* __restrict__ qw, uint16_t* __restrict__ scales,
    uint32_t* __restrict__ zeros, uint32_t* __restrict__ range_errors, int K, int g) {
    extern __shared__ uint8_t zbuf[];  // one zero-point per group of this row
    constexpr int kTeams = kQuantBlock / LPG;
    const int n = blockIdx.x;
    const int team = threadIdx.x / LPG;
    const int tl = threadIdx.x % LPG;
    const int G = K / g;
    const int wpg = g / 8;
    const float* wrow = w + (size_t)n * K;
    uint32_t* qrow = qw + (size_t)n * (K / 8);

    // every team runs the same number of rounds so that the team shuffles are
    // executed by whole waves
    const int rounds = (G + kTeams - 1) / kTeams;
    for (int r = 0; r < rounds; ++r) {
        const int grp = r * kTeams + team;
        const bool live = grp < G;
        float lo = 0.f, hi = 0.f;
        if (live) {
            for (int wi = tl; wi < wpg; wi += LPG) {
                float v[8];
                load8(wrow + (size_t)grp * g + wi * 8, v);
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    lo = fminf(lo, v[j]);
                    hi = fmaxf(hi, v[j]);
                }
            }
        }
#pragma unroll
        for (int off = 1; off < LPG; off <<= 1) {
            lo = fminf(lo, __shfl_xor(lo, off, kWave));
            hi = fmaxf(hi, __shfl_xor(hi, off, kWave));
        }
        if (!live) continue;
        float s32 = (hi - lo) / 15.0f;
        const bool over = s32 > 65504.0f;
        if (over) s32 = 65504.0f;
        uint16_t sb = f32_to_f16_bits_up(s32);
        if (sb < 0x0400) sb = 0x0400;   // 2^-14, the smallest normal fp16
        if (hi == lo) sb = 0x3C00;      // all-zero group: scale 1
        const float s = f16_bits_to_f32(sb);
        const float z = fminf(fmaxf(rintf(-lo / s), 0.f), 15.f);
        for (int wi = tl; wi < wpg; wi += LPG) {
            float v[8];
            load8(wrow + (size_t)grp * g + wi * 8, v);
            uint32_t word = 0;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float q = fminf(fmaxf(rintf(v[j] / s) + z, 0.f), 15.f);
                word |= (uint32_t)(int)q << (4 * j);
            }
            qrow[(size_t)grp * wpg + wi] = word;
        }
        if (tl == 0) {
            scales[(size_t)n * G + grp] = sb;
            zbuf[grp] = (uint8_t)(int)z;
            if (over && range_errors) atomicAdd(range_errors, 1u);
        }
    }
    __syncthreads();
    const int zwords = (G + 7) / 8;
    for (int zi = threadIdx.x; zi < zwords; zi += kQuantBlock) {
        uint32_t word = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int grp = zi * 8 + j;
            if (grp < G) word |= (uint32_t)zbuf[grp] << (4 * j);
        }
        zeros[(size_t)n * zwords + zi] = word;
    }
}

// One block per row (output channel): absmax, then codes.
__global__ __launch_bounds__(kQuantBlock) void quantize_sym_kernel(
    const float* __restrict__ w, uint32_t* __restrict__ qw, float* __restrict__ scales, int K) {
    __shared__ float red[kQuantBlock / kWave];
    const int n = blockIdx.x;
    const float* wrow = w + (size_t)n * K;
    const int words = K / 8;
    float amax = 0.f;
    for (int wi = threadIdx.x; wi < words; wi += kQuantBlock) {
        float v[8];
        load8(wrow + (size_t)wi * 8, v);
#pragma unroll
        for (int j = 0; j < 8; ++j) amax = fmaxf(amax, fabsf(v[j]));
    }
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) amax = fmaxf(amax, __shfl_xor(amax, off, kWave));
    if (threadIdx.x % kWave == 0) red[threadIdx.x / kWave] = amax;
    __syncthreads();
    amax = red[0];
#pragma unroll
    for (int i = 1; i < kQuantBlock / kWave; ++i) amax = fmaxf(amax, red[i]);
    const float s = (amax == 0.f) ? 1.0f : amax / 7.0f;
    if (threadIdx.x == 0) scales[n] = s;
    uint32_t* qrow = qw + (size_t)n * words;
    for (int wi = threadIdx.x; wi < words; wi += kQuantBlock) {
        float v[8];
        load8(wrow + (size_t)wi * 8, v);
        uint32_t word = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float q = fminf(fmaxf(rintf(v[j] / s), -8.f), 7.f);
            word |= ((uint32_t)(int)q & 0xFu) << (4 * j);
        }
        qrow[wi] = word;
    }
}

template <bool kSigned>
__global__ __launch_bounds__(256) void unpack_kernel(const uint32_t* __restrict__ qw,
                                                     uint2* __restrict__ codes, size_t words) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= words) return;
    const uint32_t w = qw[i];
    uint32_t lo = 0, hi = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        uint32_t a = (w >> (4 * j)) & 0xFu, b = (w >> (4 * (j + 4))) & 0xFu;
        if (kSigned) {
            a = (a ^ 8u) - 8u;  // sign-extend the nibble
            b = (b ^ 8u) - 8u;
        }
        lo |= (a & 0xFFu) << (8 * j);
        hi |= (b & 0xFFu) << (8 * j);
    }
    codes[i] = make_uint2(lo, hi);
}

// ---- activations ---------------------------------------------------------

__global__ void act_scale_init_kernel(float* s_a) { *reinterpret_cast<uint32_t*>(s_a) = 0u; }

// max(max(a), 0) through an integer atomic: non-negative floats are ordered
// like their bit patterns, and a tensor with no positive element leaves 0.
__global__ __launch_bounds__(256) void act_scale_reduce_kernel(const float* __restrict__ a, size_t n,
                                                               float* s_a) {
    float m = 0.f;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
        m = fmaxf(m, a[i]);
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) m = fmaxf(m, __shfl_xor(m, off, kWave));
    if (threadIdx.x % kWave == 0 && m > 0.f)
        atomicMax(reinterpret_cast<uint32_t*>(s_a), __builtin_bit_cast(uint32_t, m));
}

__global__ void act_scale_final_kernel(float* s_a) {
    const float m = *s_a;
    *s_a = (m > 0.f) ? m / 15.0f : 1.0f;
}

__global__ __launch_bounds__(256) void act_quant_kernel(const float* __restrict__ a, size_t words,
                                                        const float* __restrict__ s_a,
                                                        uint32_t* __restrict__ out) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= words) return;
    const float s = *s_a;
    float v[8];
    load8(a + i * 8, v);
    uint32_t word = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const float q = fminf(fmaxf(rintf(v[j] / s), 0.f), 15.f);
        word |= (uint32_t)(int)q << (4 * j);
    }
    out[i] = word;
}

int next_pow2(int v) {
    int p = 1;
    while (p < v) p <<= 1;
    return p;
}

}  // namespace

hipError_t launch_quantize_asym(const qail_wdesc& d, const float* w, uint32_t* qw, uint16_t* scales,
                                uint32_t* zeros, uint32_t* range_errors, hipStream_t st) {
    const int G = d.K / d.group_size;
    const size_t lds = (size_t)((G + 15) / 16) * 16;
    int lpg = next_pow2(d.group_size / 8);
    if (lpg > kWave) lpg = kWave;
    dim3 grid(d.N), block(kQuantBlock);
#define QAIL_LAUNCH_ASYM(L)                                                                          \
    case L:                                                                                          \
        hipLaunchKernelGGL(quantize_asym_kernel<L>, grid, block, lds, st, w, qw, scales, zeros,      \
                           range_errors, d.K, d.group_size);                                         \
        break;
    switch (lpg) {
        QAIL_LAUNCH_ASYM(1)
        QAIL_LAUNCH_ASYM(2)
        QAIL_LAUNCH_ASYM(4)
        QAIL_LAUNCH_ASYM(8)
        QAIL_LAUNCH_ASYM(16)
        QAIL_LAUNCH_ASYM(32)
        QAIL_LAUNCH_ASYM(64)
    }
#undef QAIL_LAUNCH_ASYM
    return hipGetLastError();
}

hipError_t launch_quantize_sym(const qail_wdesc& d, const float* w, uint32_t* qw, float* scales,
                               hipStream_t st) {
    hipLaunchKernelGGL(quantize_sym_kernel, dim3(d.N), dim3(kQuantBlock), 0, st, w, qw, scales, d.K);
    return hipGetLastError();
}

hipError_t launch_unpack(const qail_wdesc& d, const uint32_t* qw, uint8_t* codes, hipStream_t st) {
    const size_t words = (size_t)d.N * (d.K / 8);
    const unsigned blocks = (unsigned)((words + 255) / 256);
    if (d.scheme == QAIL_W4_SYM_CHANNEL)
        hipLaunchKernelGGL(unpack_kernel<true>, dim3(blocks), dim3(256), 0, st, qw,
                           reinterpret_cast<uint2*>(codes), words);
    else
        hipLaunchKernelGGL(unpack_kernel<false>, dim3(blocks), dim3(256), 0, st, qw,
                           reinterpret_cast<uint2*>(codes), words);
    return hipGetLastError();
}

hipError_t launch_act_scale(const float* a, size_t n, float* s_a, hipStream_t st) {
    hipLaunchKernelGGL(act_scale_init_kernel, dim3(1), dim3(1), 0, st, s_a);
    size_t blocks = (n + 256 * 8 - 1) / (256 * 8);
    if (blocks > 2048) blocks = 2048;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(act_scale_reduce_kernel, dim3((unsigned)blocks), dim3(256), 0, st, a, n, s_a);
    hipLaunchKernelGGL(act_scale_final_kernel, dim3(1), dim3(1), 0, st, s_a);
    return hipGetLastError();
}

hipError_t launch_act_quant(const float* a, size_t n, const float* s_a, uint32_t* out, hipStream_t st) {
    const size_t words = n / 8;
    const unsigned blocks = (unsigned)((words + 255) / 256);
    hipLaunchKernelGGL(act_quant_kernel, dim3(blocks), dim3(256), 0, st, a, words, s_a, out);
    return hipGetLastError();
}

}  // namespace qail
