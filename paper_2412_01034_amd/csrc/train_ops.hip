// Training-side operators (Sec. 4.1, Algorithm 1: the quantised policy is trained through its
// quantisers with the straight-through estimator; Sec. 4.2, Eq. 3: the QBC term, which the
// appendix instantiates as the mean L2 distance between the two policies' final logits).
// All are HBM-bound elementwise / reduction kernels.  Reductions are in a fixed order (per-block
// partial sums, then one block adds them): the results do not depend on scheduling.
#include "qail_internal.h"

namespace qail {

namespace {

constexpr int kRedBlocks = 1024;  // partial sums of the step gradient (workspace floats)

__device__ __forceinline__ float block_sum_256(float v, float* red) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, kWave);
    if (threadIdx.x % kWave == 0) red[threadIdx.x / kWave] = v;
    __syncthreads();
    const float r = (red[0] + red[1]) + (red[2] + red[3]);
    __syncthreads();
    return r;
}

// w_hat = (q - z) * s with (q, s, z) of the 4-bit group quantiser: one wave per (row, group).
__device__ __forceinline__ uint16_t f16_up(float v) {
    _Float16 h = (_Float16)v;
    uint16_t b = __builtin_bit_cast(uint16_t, h);
    if ((float)h < v) b += 1;
    return b;
}
__global__ __launch_bounds__(256) void fake_quant_w4_kernel(const float* __restrict__ w, float* __restrict__ out,
                                                            long long ngroups, int g) {
    const long long gi = (long long)blockIdx.x * 4 + threadIdx.x / kWave;
    if (gi >= ngroups) return;  // wave-uniform
    const int lane = threadIdx.x % kWave;
    const float4* src = reinterpret_cast<const float4*>(w + gi * g);
    float lo = 0.f, hi = 0.f;
    for (int i = lane; i < g / 4; i += kWave) {
        const float4 v = src[i];
        lo = fminf(fminf(lo, fminf(v.x, v.y)), fminf(v.z, v.w));
        hi = fmaxf(fmaxf(hi, fmaxf(v.x, v.y)), fmaxf(v.z, v.w));
    }
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        lo = fminf(lo, __shfl_xor(lo, o, kWave));
        hi = fmaxf(hi, __shfl_xor(hi, o, kWave));
    }
    float s32 = (hi - lo) / 15.0f;
    if (s32 > 65504.0f) s32 = 65504.0f;
    uint16_t sb = f16_up(s32);
    if (sb < 0x0400) sb = 0x0400;
    if (hi == lo) sb = 0x3C00;
    const float s = f16_bits_to_f32(sb);
    const float z = fminf(fmaxf(rintf(-lo / s), 0.f), 15.f);
    float4* dst = reinterpret_cast<float4*>(out + gi * g);
    for (int i = lane; i < g / 4; i += kWave) {
        const float4 v = src[i];
        float4 r;
        r.x = (fminf(fmaxf(rintf(v.x / s) + z, 0.f), 15.f) - z) * s;
        r.y = (fminf(fmaxf(rintf(v.y / s) + z, 0.f), 15.f) - z) * s;
        r.z = (fminf(fmaxf(rintf(v.z / s) + z, 0.f), 15.f) - z) * s;
        r.w = (fminf(fmaxf(rintf(v.w / s) + z, 0.f), 15.f) - z) * s;
        dst[i] = r;
    }
}

// The same for groups of at most 128 * kPer values: half a wave per group, the group held in
// registers (read once), a block walks over groups 8 at a time.
template <int kPer>
__global__ __launch_bounds__(256) void fake_quant_w4_half_kernel(const float* __restrict__ w, float* __restrict__ out,
                                                                 long long ngroups, int g) {
    const int half = threadIdx.x / 32, l = threadIdx.x % 32;
    const int n4 = g / 4;
    for (long long gi = (long long)blockIdx.x * 8 + half; gi < ngroups; gi += (long long)gridDim.x * 8) {
        const float4* src = reinterpret_cast<const float4*>(w + gi * g);
        float4 v[kPer];
        float lo = 0.f, hi = 0.f;
#pragma unroll
        for (int u = 0; u < kPer; ++u) {
            v[u] = l + 32 * u < n4 ? src[l + 32 * u] : make_float4(0.f, 0.f, 0.f, 0.f);  // 0 leaves lo <= 0 <= hi alone
            lo = fminf(fminf(lo, fminf(v[u].x, v[u].y)), fminf(v[u].z, v[u].w));
            hi = fmaxf(fmaxf(hi, fmaxf(v[u].x, v[u].y)), fmaxf(v[u].z, v[u].w));
        }
#pragma unroll
        for (int o = 1; o < 32; o <<= 1) {
            lo = fminf(lo, __shfl_xor(lo, o, kWave));
            hi = fmaxf(hi, __shfl_xor(hi, o, kWave));
        }
        float s32 = (hi - lo) / 15.0f;
        if (s32 > 65504.0f) s32 = 65504.0f;
        uint16_t sb = f16_up(s32);
        if (sb < 0x0400) sb = 0x0400;
        if (hi == lo) sb = 0x3C00;
        const float s = f16_bits_to_f32(sb);
        const float z = fminf(fmaxf(rintf(-lo / s), 0.f), 15.f);
        float4* dst = reinterpret_cast<float4*>(out + gi * g);
#pragma unroll
        for (int u = 0; u < kPer; ++u) {
            float4 r;
            r.x = (fminf(fmaxf(rintf(v[u].x / s) + z, 0.f), 15.f) - z) * s;
            r.y = (fminf(fmaxf(rintf(v[u].y / s) + z, 0.f), 15.f) - z) * s;
            r.z = (fminf(fmaxf(rintf(v[u].z / s) + z, 0.f), 15.f) - z) * s;
            r.w = (fminf(fmaxf(rintf(v[u].w / s) + z, 0.f), 15.f) - z) * s;
            if (l + 32 * u < n4) dst[l + 32 * u] = r;
        }
    }
}

// Four values per thread and access (the arrays are 16-byte aligned); the last n % 4 values one by one.
__global__ __launch_bounds__(256) void lsq_fwd_kernel(const float* __restrict__ v, size_t n, const float* __restrict__ sp,
                                                      float qn, float qp, float* __restrict__ out) {
    const float s = *sp;
    const size_t n4 = n / 4, stride = (size_t)gridDim.x * 256, first = (size_t)blockIdx.x * 256 + threadIdx.x;
    const float4* v4 = reinterpret_cast<const float4*>(v);
    float4* o4 = reinterpret_cast<float4*>(out);
    for (size_t i = first; i < n4; i += stride) {
        const float4 a = v4[i];
        float4 r;
        r.x = fminf(fmaxf(rintf(a.x / s), qn), qp) * s;
        r.y = fminf(fmaxf(rintf(a.y / s), qn), qp) * s;
        r.z = fminf(fmaxf(rintf(a.z / s), qn), qp) * s;
        r.w = fminf(fmaxf(rintf(a.w / s), qn), qp) * s;
        o4[i] = r;
    }
    for (size_t i = n4 * 4 + first; i < n; i += stride) out[i] = fminf(fmaxf(rintf(v[i] / s), qn), qp) * s;
}

__global__ __launch_bounds__(256) void lsq_bwd_kernel(const float* __restrict__ v, const float* __restrict__ dout, size_t n,
                                                      const float* __restrict__ sp, float qn, float qp,
                                                      float* __restrict__ dv, float* __restrict__ partial) {
    __shared__ float red[4];
    const float s = *sp;
    float acc = 0.f;
    auto one = [&](float vi, float d, float& g) {
        const float r = vi / s;
        const bool inside = r >= qn && r <= qp;
        g = inside ? d : 0.f;
        const float t = inside ? rintf(r) - r : (r < qn ? qn : qp);
        acc = fmaf(d, t, acc);
    };
    const size_t n4 = n / 4, stride = (size_t)gridDim.x * 256, first = (size_t)blockIdx.x * 256 + threadIdx.x;
    const float4* v4 = reinterpret_cast<const float4*>(v);
    const float4* d4 = reinterpret_cast<const float4*>(dout);
    float4* g4 = reinterpret_cast<float4*>(dv);
    for (size_t i = first; i < n4; i += stride) {
        const float4 a = v4[i], d = d4[i];
        float4 g;
        one(a.x, d.x, g.x);
        one(a.y, d.y, g.y);
        one(a.z, d.z, g.z);
        one(a.w, d.w, g.w);
        g4[i] = g;
    }
    for (size_t i = n4 * 4 + first; i < n; i += stride) one(v[i], dout[i], dv[i]);
    const float tot = block_sum_256(acc, red);
    if (threadIdx.x == 0) partial[blockIdx.x] = tot;
}

__global__ __launch_bounds__(256) void sum_partials_kernel(const float* __restrict__ partial, int count, float mul,
                                                           float* __restrict__ out) {
    __shared__ float red[4];
    float acc = 0.f;
    for (int i = threadIdx.x; i < count; i += 256) acc += partial[i];
    const float tot = block_sum_256(acc, red);
    if (threadIdx.x == 0) *out = mul * tot;
}

// One block per batch row: distance, then (optionally) the row of the gradient.
__global__ __launch_bounds__(256) void qbc_rows_kernel(const float* __restrict__ lq, const float* __restrict__ lf, int D,
                                                       float inv_b, float* __restrict__ dist, float* __restrict__ grad) {
    __shared__ float red[4];
    const size_t base = (size_t)blockIdx.x * D;
    float acc = 0.f;
    for (int j = threadIdx.x; j < D; j += 256) {
        const float d = lq[base + j] - lf[base + j];
        acc = fmaf(d, d, acc);
    }
    const float nrm = sqrtf(block_sum_256(acc, red));
    if (threadIdx.x == 0) dist[blockIdx.x] = nrm;
    if (grad) {
        const float k = nrm > 0.f ? inv_b / nrm : 0.f;
        for (int j = threadIdx.x; j < D; j += 256) grad[base + j] = (lq[base + j] - lf[base + j]) * k;
    }
}

// The same with 1024 threads per row and the row's differences held in registers (D a multiple
// of 4, at most 32768): the logits are read once.
constexpr int kQbcPer = 8;   // 16-byte pieces per thread
__global__ __launch_bounds__(1024) void qbc_rows_reg_kernel(const float* __restrict__ lq, const float* __restrict__ lf, int D,
                                                            float inv_b, float* __restrict__ dist, float* __restrict__ grad) {
    __shared__ float red[16];
    const size_t base4 = (size_t)blockIdx.x * (D / 4);
    const float4* q4 = reinterpret_cast<const float4*>(lq) + base4;
    const float4* f4 = reinterpret_cast<const float4*>(lf) + base4;
    const int n4 = D / 4;
    float4 d[kQbcPer];
    float acc = 0.f;
#pragma unroll
    for (int u = 0; u < kQbcPer; ++u) {
        const int j = threadIdx.x + 1024 * u;
        d[u] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (j < n4) {
            const float4 a = q4[j], b = f4[j];
            d[u] = make_float4(a.x - b.x, a.y - b.y, a.z - b.z, a.w - b.w);
        }
        acc = fmaf(d[u].x, d[u].x, acc);
        acc = fmaf(d[u].y, d[u].y, acc);
        acc = fmaf(d[u].z, d[u].z, acc);
        acc = fmaf(d[u].w, d[u].w, acc);
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) acc += __shfl_xor(acc, o, kWave);
    if (threadIdx.x % kWave == 0) red[threadIdx.x / kWave] = acc;
    __syncthreads();
    float tot = 0.f;
#pragma unroll
    for (int w = 0; w < 16; ++w) tot += red[w];
    const float nrm = sqrtf(tot);
    if (threadIdx.x == 0) dist[blockIdx.x] = nrm;
    if (grad) {
        const float k = nrm > 0.f ? inv_b / nrm : 0.f;
        float4* g4 = reinterpret_cast<float4*>(grad) + base4;
#pragma unroll
        for (int u = 0; u < kQbcPer; ++u) {
            const int j = threadIdx.x + 1024 * u;
            if (j < n4) g4[j] = make_float4(d[u].x * k, d[u].y * k, d[u].z * k, d[u].w * k);
        }
    }
}

}  // namespace

hipError_t launch_fake_quant_w4(const qail_wdesc& d, const float* w, float* out, hipStream_t st) {
    const long long ngroups = (long long)d.N * (d.K / d.group_size);
    if (d.group_size <= 256) {
        long long blocks = (ngroups + 7) / 8;
        if (blocks > 4096) blocks = 4096;
        if (d.group_size <= 128)
            hipLaunchKernelGGL(fake_quant_w4_half_kernel<1>, dim3((unsigned)blocks), dim3(256), 0, st, w, out, ngroups, d.group_size);
        else
            hipLaunchKernelGGL(fake_quant_w4_half_kernel<2>, dim3((unsigned)blocks), dim3(256), 0, st, w, out, ngroups, d.group_size);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(fake_quant_w4_kernel, dim3((unsigned)((ngroups + 3) / 4)), dim3(256), 0, st, w, out, ngroups,
                       d.group_size);
    return hipGetLastError();
}

hipError_t launch_lsq_fwd(const float* v, size_t n, const float* s, int qn, int qp, float* out, hipStream_t st) {
    size_t blocks = (n / 4 + 255) / 256 + 1;
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(lsq_fwd_kernel, dim3((unsigned)blocks), dim3(256), 0, st, v, n, s, (float)qn, (float)qp, out);
    return hipGetLastError();
}

size_t lsq_bwd_workspace() { return kRedBlocks * sizeof(float); }

hipError_t launch_lsq_bwd(const float* v, const float* dout, size_t n, const float* s, int qn, int qp, float grad_scale,
                          float* dv, float* ds, float* ws, hipStream_t st) {
    size_t blocks = (n / 4 + 255) / 256 + 1;
    if (blocks > kRedBlocks) blocks = kRedBlocks;
    hipLaunchKernelGGL(lsq_bwd_kernel, dim3((unsigned)blocks), dim3(256), 0, st, v, dout, n, s, (float)qn, (float)qp, dv, ws);
    hipLaunchKernelGGL(sum_partials_kernel, dim3(1), dim3(256), 0, st, ws, (int)blocks, grad_scale, ds);
    return hipGetLastError();
}

hipError_t launch_qbc(const float* lq, const float* lf, int B, int D, float* loss, float* grad, float* ws, hipStream_t st) {
    const bool aligned = ((reinterpret_cast<uintptr_t>(lq) | reinterpret_cast<uintptr_t>(lf) | reinterpret_cast<uintptr_t>(grad)) & 15u) == 0;
    if (D % 4 == 0 && D <= 1024 * 4 * kQbcPer && aligned)
        hipLaunchKernelGGL(qbc_rows_reg_kernel, dim3(B), dim3(1024), 0, st, lq, lf, D, 1.0f / (float)B, ws, grad);
    else
        hipLaunchKernelGGL(qbc_rows_kernel, dim3(B), dim3(256), 0, st, lq, lf, D, 1.0f / (float)B, ws, grad);
    hipLaunchKernelGGL(sum_partials_kernel, dim3(1), dim3(256), 0, st, ws, B, 1.0f / (float)B, loss);
    return hipGetLastError();
}

}  // namespace qail
